// Winograd F(m x m, 3 x 3) transform matrices used by the GPU kernels.
//
// The paper names the Winograd kernel family (Table 2, Fig. 3) without printing
// matrices; these are the Toom-Cook interpolation matrices for
//   set 0 (F2)  : points 0, 1, -1                     (4x4 tiles)
//   set 1 (F4)  : points 0, 1, -1, 2, -2              (6x6 tiles, float32 storage)
//   set 2 (F4H) : points 0, 1, -1, 2, -1/2, with G rows scaled by 4,4,4,16,4,1 and
//                 the columns of A^T divided by the same factors (6x6 tiles, float16
//                 storage: smaller spread of U, smaller entries in A^T)
//   set 3 (F6)  : points 0, 1, -1, 2, -2, 1/2, -1/2   (8x8 tiles, float32 storage)
// written out literally.  G is alpha x 3, BT is alpha x alpha, AT is m x alpha.
#pragma once

namespace nnv {

template <int SET> struct WinoMat;

template <> struct WinoMat<0> {
    static constexpr int M = 2, A = 4;
    static constexpr float G[4][3] = {{1.f, 0.f, 0.f}, {.5f, .5f, .5f}, {.5f, -.5f, .5f}, {0.f, 0.f, 1.f}};
    static constexpr float BT[4][4] = {{1, 0, -1, 0}, {0, 1, 1, 0}, {0, -1, 1, 0}, {0, 1, 0, -1}};
    static constexpr float AT[2][4] = {{1, 1, 1, 0}, {0, 1, -1, -1}};
};

template <> struct WinoMat<1> {
    static constexpr int M = 4, A = 6;
    static constexpr float G[6][3] = {{1.f / 4, 0.f, 0.f},
                                      {-1.f / 6, -1.f / 6, -1.f / 6},
                                      {-1.f / 6, 1.f / 6, -1.f / 6},
                                      {1.f / 24, 1.f / 12, 1.f / 6},
                                      {1.f / 24, -1.f / 12, 1.f / 6},
                                      {0.f, 0.f, 1.f}};
    static constexpr float BT[6][6] = {{4, 0, -5, 0, 1, 0},  {0, -4, -4, 1, 1, 0}, {0, 4, -4, -1, 1, 0},
                                       {0, -2, -1, 2, 1, 0}, {0, 2, -1, -2, 1, 0}, {0, 4, 0, -5, 0, 1}};
    static constexpr float AT[4][6] = {{1, 1, 1, 1, 1, 0}, {0, 1, -1, 2, -2, 0}, {0, 1, 1, 4, 4, 0}, {0, 1, -1, 8, -8, 1}};
};

template <> struct WinoMat<2> {
    static constexpr int M = 4, A = 6;
    static constexpr float G[6][3] = {{4.f, 0.f, 0.f},
                                      {-4.f / 3, -4.f / 3, -4.f / 3},
                                      {4.f / 3, -4.f / 3, 4.f / 3},
                                      {16.f / 15, 32.f / 15, 64.f / 15},
                                      {-64.f / 15, 32.f / 15, -16.f / 15},
                                      {0.f, 0.f, 1.f}};
    static constexpr float BT[6][6] = {{1, 1.5f, -2, -1.5f, 1, 0},  {0, -1, -2.5f, -.5f, 1, 0}, {0, 1, .5f, -2.5f, 1, 0},
                                       {0, -.5f, -1, .5f, 1, 0},    {0, 2, -1, -2, 1, 0},       {0, 1, 1.5f, -2, -1.5f, 1}};
    static constexpr float AT[4][6] = {{.25f, .25f, .25f, .0625f, .25f, 0},
                                       {0, .25f, -.25f, .125f, -.125f, 0},
                                       {0, .25f, .25f, .25f, .0625f, 0},
                                       {0, .25f, -.25f, .5f, -.03125f, 1}};
};

template <> struct WinoMat<3> {
    static constexpr int M = 6, A = 8;
    static constexpr float G[8][3] = {{1.f, 0.f, 0.f},
                                      {-2.f / 9, -2.f / 9, -2.f / 9},
                                      {-2.f / 9, 2.f / 9, -2.f / 9},
                                      {1.f / 90, 1.f / 45, 2.f / 45},
                                      {1.f / 90, -1.f / 45, 2.f / 45},
                                      {32.f / 45, 16.f / 45, 8.f / 45},
                                      {32.f / 45, -16.f / 45, 8.f / 45},
                                      {0.f, 0.f, 1.f}};
    static constexpr float BT[8][8] = {{1, 0, -5.25f, 0, 5.25f, 0, -1, 0},
                                       {0, 1, 1, -4.25f, -4.25f, 1, 1, 0},
                                       {0, -1, 1, 4.25f, -4.25f, -1, 1, 0},
                                       {0, .5f, .25f, -2.5f, -1.25f, 2, 1, 0},
                                       {0, -.5f, .25f, 2.5f, -1.25f, -2, 1, 0},
                                       {0, 2, 4, -2.5f, -5, .5f, 1, 0},
                                       {0, -2, 4, 2.5f, -5, -.5f, 1, 0},
                                       {0, -1, 0, 5.25f, 0, -5.25f, 0, 1}};
    static constexpr float AT[6][8] = {{1, 1, 1, 1, 1, 1, 1, 0},
                                       {0, 1, -1, 2, -2, .5f, -.5f, 0},
                                       {0, 1, 1, 4, 4, .25f, .25f, 0},
                                       {0, 1, -1, 8, -8, .125f, -.125f, 0},
                                       {0, 1, 1, 16, 16, .0625f, .0625f, 0},
                                       {0, 1, -1, 32, -32, .03125f, -.03125f, 1}};
};

}  // namespace nnv
