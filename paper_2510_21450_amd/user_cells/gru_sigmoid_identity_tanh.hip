// Example of a cell added from outside the library: the diagonal GRU (Eq. (7a),
// Eq. (9)) with the reset nonlinearity replaced by the identity (App. D.3 makes
// the nonlinearities parameters of the cell): the candidate reads
// a_c (a_r h + u_r + b_r) h, a quadratic in the previous state, inside tanh.
// Exports gru_sigmoid_identity_tanh_forward / _backward / ...
#include "pararnn_cell.h"
#include "pararnn_nonlin.h"

using GruSigmoidIdentityTanh = pararnn::GruDiagNl<pararnn::NlSigmoid, pararnn::NlIdentity, pararnn::NlTanh>;
PARARNN_DEFINE_CELL(GruSigmoidIdentityTanh, gru_sigmoid_identity_tanh)
