// Example of a cell added from outside the library: the diagonal GRU (Eq. (7a),
// Eq. (9)) with a softsign reset gate and no state nonlinearity (App. D.3 makes
// the nonlinearities parameters of the cell): the candidate is linear in its
// input, c = a_c (r h) + u_c + b_c, so the state is not confined to (-1, 1).
// Exports gru_sigmoid_softsign_identity_forward / _backward / ...
#include "pararnn_cell.h"
#include "pararnn_nonlin.h"

using GruSigmoidSoftsignIdentity = pararnn::GruDiagNl<pararnn::NlSigmoid, pararnn::NlSoftsign, pararnn::NlIdentity>;
PARARNN_DEFINE_CELL(GruSigmoidSoftsignIdentity, gru_sigmoid_softsign_identity)
