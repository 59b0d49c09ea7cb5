// Example of a cell added from outside the library: the diagonal GRU (Eq. (7a),
// Eq. (9)) with the state nonlinearity replaced by softsign, built from the
// selectable-nonlinearity template.  Exports gru_softsign_forward / _backward / ...
#include "pararnn_cell.h"
#include "pararnn_nonlin.h"

using GruSoftsign = pararnn::GruDiagNl<pararnn::NlSigmoid, pararnn::NlSigmoid, pararnn::NlSoftsign>;
PARARNN_DEFINE_CELL(GruSoftsign, gru_softsign)
