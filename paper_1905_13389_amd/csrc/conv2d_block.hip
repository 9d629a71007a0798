// The convolution kernels of conv2d_tile.h with the residual-block terms (bias, shortcut) compiled
// into the epilogue; qnn_conv2d_block launches these when it is given any such term.
#include "conv2d_tile.h"

namespace qnn {

int conv_tiles_block(int wb, int ab, const ConvTileParams &p, hipStream_t st) { return conv_dispatch<true>(wb, ab, p, st); }

} // namespace qnn
