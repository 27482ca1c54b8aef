// Instantiations of the implicit-GEMM convolution kernel for the rectangular and
// 5x5 filters of Inception-style networks (1x7, 7x1, 1x3, 3x1, 5x5), forward and,
// through the stride-1 duality of Section II-I, backward by data.  The kernel is
// the one the square ResNet filters use; only the compile-time filter extent and
// the per-thread share of the staged input tile differ.
#include "igemm_kernel.h"

namespace convmi {

// The wave layouts the planner tries, each with two and three staged positions
// per thread (the tiles of 8x8 to 35x35 images need no more).
#define RECT_F32(R, S)                                   \
    IGEMM_ENTRY(CONV_F32, 4, 1, 1, 7, 2, R, S, 2),       \
    IGEMM_ENTRY(CONV_F32, 4, 1, 1, 7, 2, R, S, 3),       \
    IGEMM_ENTRY(CONV_F32, 2, 2, 1, 7, 2, R, S, 2),       \
    IGEMM_ENTRY(CONV_F32, 2, 2, 1, 7, 2, R, S, 3),       \
    IGEMM_ENTRY(CONV_F32, 2, 2, 1, 7, 1, R, S, 3)
#define RECT_BF16(R, S)                                  \
    IGEMM_ENTRY(CONV_BF16, 1, 4, 2, 4, 2, R, S, 2),      \
    IGEMM_ENTRY(CONV_BF16, 1, 4, 2, 4, 2, R, S, 3),      \
    IGEMM_ENTRY(CONV_BF16, 2, 2, 2, 7, 2, R, S, 2),      \
    IGEMM_ENTRY(CONV_BF16, 2, 2, 2, 7, 2, R, S, 3),      \
    IGEMM_ENTRY(CONV_BF16, 2, 2, 1, 7, 1, R, S, 3)

static IgemmEntry g_rect[] = {
    RECT_F32(1, 7), RECT_F32(7, 1), RECT_F32(1, 3), RECT_F32(3, 1),
    RECT_BF16(1, 7), RECT_BF16(7, 1), RECT_BF16(1, 3), RECT_BF16(3, 1),
    // 5x5: 25 taps of weights per channel block; one channel block per step keeps two
    // buffers of a 128-row weight tile within the LDS
    IGEMM_ENTRY(CONV_F32, 2, 2, 1, 7, 1, 5, 5, 3),
    IGEMM_ENTRY(CONV_F32, 2, 2, 1, 7, 2, 5, 5, 3),
    IGEMM_ENTRY(CONV_F32, 4, 1, 1, 7, 1, 5, 5, 3),
    IGEMM_ENTRY(CONV_BF16, 1, 4, 2, 4, 2, 5, 5, 3),
    IGEMM_ENTRY(CONV_BF16, 1, 4, 2, 4, 1, 5, 5, 3),
    IGEMM_ENTRY(CONV_BF16, 2, 2, 1, 7, 1, 5, 5, 3),
    // strided 3x3 over an image with a single channel block and rows as wide as the tile
    // (the first layer of a 299 x 299 network): four staged positions per thread
    IGEMM_ENTRY(CONV_F32, 2, 2, 1, 7, 1, 3, 3, 4),
    IGEMM_ENTRY(CONV_BF16, 2, 2, 1, 7, 1, 3, 3, 4),
    // strided 3x3 of the grid-reduction modules: the input tile of a full pixel tile
    // spans twice its rows and columns
    IGEMM_ENTRY(CONV_F32, 4, 1, 1, 7, 2, 3, 3, 4),
    IGEMM_ENTRY(CONV_F32, 2, 2, 1, 7, 2, 3, 3, 4),
    IGEMM_ENTRY(CONV_BF16, 4, 1, 1, 7, 2, 3, 3, 4),
    // 3x3 results with at most 32 channel rows (the 32-channel stem layers and their
    // backward passes): 32 rows x 896 pixels per workgroup
    IGEMM_ENTRY(CONV_F32, 1, 4, 1, 7, 2, 3, 3, 5),
    IGEMM_ENTRY(CONV_F32, 1, 4, 1, 7, 2, 3, 3, 3),
    // (six rows of a 147-wide image fill the pixel slots; a band that crosses two images
    // spans ten input rows)
    IGEMM_ENTRY(CONV_F32, 1, 4, 1, 7, 2, 3, 3, 6),
    IGEMM_ENTRY(CONV_BF16, 1, 4, 1, 7, 2, 3, 3, 6),
    // ... with a single input channel block under stride 2 (the 3-channel first layer of a
    // 299 x 299 network: six 149-pixel output rows fill the 896 pixel slots, their input tile
    // is 13 rows of 299), and the 2x2 residue classes of that layer's backward pass
    IGEMM_ENTRY(CONV_F32, 1, 4, 1, 7, 1, 3, 3, 16),
    IGEMM_ENTRY(CONV_BF16, 1, 4, 1, 7, 1, 3, 3, 16),
    IGEMM_ENTRY(CONV_F32, 1, 4, 1, 7, 2, 2, 2, 4),
    IGEMM_ENTRY(CONV_F32, 1, 4, 1, 7, 2, 2, 2, 5),
};

IgemmEntry *igemm_rect_entries(int *count)
{
    *count = (int)(sizeof(g_rect) / sizeof(g_rect[0]));
    return g_rect;
}

}  // namespace convmi
