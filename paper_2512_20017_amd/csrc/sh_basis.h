// Real spherical-harmonics basis to degree 3 and its gradient: the view-dependent colour of a point is
// max(0, 0.5 + sum_k Y_k(dir) sh_k) (a reading of "view-dependent color", paper Sec. 2.1). Shared by the 3D-Gaussian and
// the 2D-surfel preprocessing kernels.
#pragma once
#include <hip/hip_runtime.h>

namespace pbdr {

// Real SH basis, index l*l+l+m, Condon-Shortley phase kept (so l=1 is (-y, z, -x)).
__device__ __forceinline__ void sh_basis(int deg, float x, float y, float z, float Y[16])
{
    Y[0] = 0.28209479177387814f;
    if (deg < 1) return;
    Y[1] = -0.4886025119029199f * y; Y[2] = 0.4886025119029199f * z; Y[3] = -0.4886025119029199f * x;
    if (deg < 2) return;
    const float xx = x * x, yy = y * y, zz = z * z;
    Y[4] = 1.0925484305920792f * x * y;
    Y[5] = -1.0925484305920792f * y * z;
    Y[6] = 0.31539156525252005f * (2.f * zz - xx - yy);
    Y[7] = -1.0925484305920792f * x * z;
    Y[8] = 0.5462742152960396f * (xx - yy);
    if (deg < 3) return;
    Y[9] = -0.5900435899266435f * y * (3.f * xx - yy);
    Y[10] = 2.890611442640554f * x * y * z;
    Y[11] = -0.4570457994644658f * y * (4.f * zz - xx - yy);
    Y[12] = 0.3731763325901154f * z * (2.f * zz - 3.f * xx - 3.f * yy);
    Y[13] = -0.4570457994644658f * x * (4.f * zz - xx - yy);
    Y[14] = 1.445305721320277f * z * (xx - yy);
    Y[15] = -0.5900435899266435f * x * (xx - 3.f * yy);
}

// d(colour)/d(direction): partial derivatives of the SH polynomials contracted with the coefficients.
__device__ __forceinline__ void sh_basis_grad(int deg, float x, float y, float z, float dY[16][3])
{
#pragma unroll
    for (int k = 0; k < 16; ++k) dY[k][0] = dY[k][1] = dY[k][2] = 0.f;
    if (deg < 1) return;
    const float c1 = 0.4886025119029199f;
    dY[1][1] = -c1; dY[2][2] = c1; dY[3][0] = -c1;
    if (deg < 2) return;
    const float c2a = 1.0925484305920792f, c2b = 0.31539156525252005f, c2c = 0.5462742152960396f;
    dY[4][0] = c2a * y; dY[4][1] = c2a * x;
    dY[5][1] = -c2a * z; dY[5][2] = -c2a * y;
    dY[6][0] = -2.f * c2b * x; dY[6][1] = -2.f * c2b * y; dY[6][2] = 4.f * c2b * z;
    dY[7][0] = -c2a * z; dY[7][2] = -c2a * x;
    dY[8][0] = 2.f * c2c * x; dY[8][1] = -2.f * c2c * y;
    if (deg < 3) return;
    const float c3a = 0.5900435899266435f, c3b = 2.890611442640554f, c3c = 0.4570457994644658f,
                c3d = 0.3731763325901154f, c3e = 1.445305721320277f;
    const float xx = x * x, yy = y * y, zz = z * z;
    dY[9][0] = -6.f * c3a * x * y;             dY[9][1] = -3.f * c3a * (xx - yy);
    dY[10][0] = c3b * y * z;                   dY[10][1] = c3b * x * z;                  dY[10][2] = c3b * x * y;
    dY[11][0] = 2.f * c3c * x * y;             dY[11][1] = -c3c * (4.f * zz - xx - 3.f * yy); dY[11][2] = -8.f * c3c * y * z;
    dY[12][0] = -6.f * c3d * x * z;            dY[12][1] = -6.f * c3d * y * z;           dY[12][2] = 3.f * c3d * (2.f * zz - xx - yy);
    dY[13][0] = -c3c * (4.f * zz - 3.f * xx - yy); dY[13][1] = 2.f * c3c * x * y;        dY[13][2] = -8.f * c3c * x * z;
    dY[14][0] = 2.f * c3e * x * z;             dY[14][1] = -2.f * c3e * y * z;           dY[14][2] = c3e * (xx - yy);
    dY[15][0] = -3.f * c3a * (xx - yy);        dY[15][1] = 6.f * c3a * x * y;
}

}  // namespace pbdr
