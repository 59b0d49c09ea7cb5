// Example of a cell added from outside the library: the diagonal GRU (Eq. (7a),
// Eq. (9)) with a tanh reset gate (range (-1, 1): it can flip the sign of the
// state the candidate reads) and a softsign state nonlinearity (App. D.3 makes
// the nonlinearities parameters of the cell).
// Exports gru_sigmoid_tanh_softsign_forward / _backward / ...
#include "pararnn_cell.h"
#include "pararnn_nonlin.h"

using GruSigmoidTanhSoftsign = pararnn::GruDiagNl<pararnn::NlSigmoid, pararnn::NlTanh, pararnn::NlSoftsign>;
PARARNN_DEFINE_CELL(GruSigmoidTanhSoftsign, gru_sigmoid_tanh_softsign)
