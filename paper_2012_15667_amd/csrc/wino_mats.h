// Transform matrices of Winograd F(m x m, 3 x 3) for m = 2, 3, 4, 6 (Sec. 2.3), in the paper's naming:
// input transform V = B d B^T, kernel transform U = L g L^T, output transform Y = A M A^T.
// They are the published Toom-Cook matrices for the interpolation points
//   m = 2: {0, 1, -1, inf}            m = 3: {0, 1, -1, 2, inf}
//   m = 4: {0, 1, -1, 2, -2, inf}     m = 6: {0, 1, -1, 2, -2, 1/2, -1/2, inf}
// and satisfy, for every output i < m, tap j < 3 and input k < m + 2:
//   sum_xi A[i][xi] * L[xi][j] * B[xi][k] = (k == i + j).
#ifndef IOLB_WINO_MATS_H
#define IOLB_WINO_MATS_H

namespace iolb {

template <int M> struct Mats;

template <> struct Mats<2> {
    static constexpr int n = 4;
    static constexpr float B[4][4] = {{1, 0, -1, 0}, {0, 1, 1, 0}, {0, -1, 1, 0}, {0, 1, 0, -1}};
    static constexpr float L[4][3] = {{1, 0, 0}, {0.5f, 0.5f, 0.5f}, {0.5f, -0.5f, 0.5f}, {0, 0, 1}};
    static constexpr float A[2][4] = {{1, 1, 1, 0}, {0, 1, -1, -1}};
};
template <> struct Mats<3> {
    static constexpr int n = 5;
    static constexpr float B[5][5] = {{2, -1, -2, 1, 0}, {0, -2, -1, 1, 0}, {0, 2, -3, 1, 0}, {0, -1, 0, 1, 0}, {0, 2, -1, -2, 1}};
    static constexpr float L[5][3] = {{1.f / 2, 0, 0},
                                      {-1.f / 2, -1.f / 2, -1.f / 2},
                                      {-1.f / 6, 1.f / 6, -1.f / 6},
                                      {1.f / 6, 1.f / 3, 2.f / 3},
                                      {0, 0, 1}};
    static constexpr float A[3][5] = {{1, 1, 1, 1, 0}, {0, 1, -1, 2, 0}, {0, 1, 1, 4, 1}};
};
template <> struct Mats<4> {
    static constexpr int n = 6;
    static constexpr float B[6][6] = {{4, 0, -5, 0, 1, 0},  {0, -4, -4, 1, 1, 0}, {0, 4, -4, -1, 1, 0},
                                      {0, -2, -1, 2, 1, 0}, {0, 2, -1, -2, 1, 0}, {0, 4, 0, -5, 0, 1}};
    static constexpr float L[6][3] = {{1.f / 4, 0, 0},
                                      {-1.f / 6, -1.f / 6, -1.f / 6},
                                      {-1.f / 6, 1.f / 6, -1.f / 6},
                                      {1.f / 24, 1.f / 12, 1.f / 6},
                                      {1.f / 24, -1.f / 12, 1.f / 6},
                                      {0, 0, 1}};
    static constexpr float A[4][6] = {{1, 1, 1, 1, 1, 0}, {0, 1, -1, 2, -2, 0}, {0, 1, 1, 4, 4, 0}, {0, 1, -1, 8, -8, 1}};
};
template <> struct Mats<6> {
    static constexpr int n = 8;
    static constexpr float B[8][8] = {{1, 0, -5.25f, 0, 5.25f, 0, -1, 0},
                                      {0, 1, 1, -4.25f, -4.25f, 1, 1, 0},
                                      {0, -1, 1, 4.25f, -4.25f, -1, 1, 0},
                                      {0, 0.5f, 0.25f, -2.5f, -1.25f, 2, 1, 0},
                                      {0, -0.5f, 0.25f, 2.5f, -1.25f, -2, 1, 0},
                                      {0, 2, 4, -2.5f, -5, 0.5f, 1, 0},
                                      {0, -2, 4, 2.5f, -5, -0.5f, 1, 0},
                                      {0, -1, 0, 5.25f, 0, -5.25f, 0, 1}};
    static constexpr float L[8][3] = {{1, 0, 0},
                                      {-2.f / 9, -2.f / 9, -2.f / 9},
                                      {-2.f / 9, 2.f / 9, -2.f / 9},
                                      {1.f / 90, 1.f / 45, 2.f / 45},
                                      {1.f / 90, -1.f / 45, 2.f / 45},
                                      {32.f / 45, 16.f / 45, 8.f / 45},
                                      {32.f / 45, -16.f / 45, 8.f / 45},
                                      {0, 0, 1}};
    static constexpr float A[6][8] = {{1, 1, 1, 1, 1, 1, 1, 0},
                                      {0, 1, -1, 2, -2, 0.5f, -0.5f, 0},
                                      {0, 1, 1, 4, 4, 0.25f, 0.25f, 0},
                                      {0, 1, -1, 8, -8, 0.125f, -0.125f, 0},
                                      {0, 1, 1, 16, 16, 0.0625f, 0.0625f, 0},
                                      {0, 1, -1, 32, -32, 0.03125f, -0.03125f, 1}};
};

}  // namespace iolb

#endif
