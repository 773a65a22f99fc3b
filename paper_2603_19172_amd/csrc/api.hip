// Context, error text, workspace size and the host-side depth schedule.
#include <math.h>
#include <new>

#include "common.hpp"
#include "ffn_layout.hpp"

extern "C" {

int dymoe_create(dymoe_ctx** out, int device)
{
    DYMOE_REQUIRE(out != nullptr && device >= 0);
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || device >= n) return DYMOE_EHIP;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return DYMOE_EHIP;
    dymoe_ctx* c = new (std::nothrow) dymoe_ctx;
    if (!c) return DYMOE_EHIP;
    c->device = device;
    c->num_cu = prop.multiProcessorCount;
    *out = c;
    return DYMOE_OK;
}

void dymoe_destroy(dymoe_ctx* ctx) { delete ctx; }

const char* dymoe_strerror(int code)
{
    switch (code) {
    case DYMOE_OK: return "success";
    case DYMOE_EINVAL: return "invalid argument";
    case DYMOE_ENOSPC: return "workspace too small";
    case DYMOE_EHIP: return "HIP runtime call failed";
    case DYMOE_ENOTSUP: return "size or mode not supported by the kernels";
    case DYMOE_ENOCTX: return "context is NULL";
    default: return "unknown error code";
    }
}

size_t dymoe_workspace_bytes(int T, int H, int F, int E, int k)
{
    if (T < 0 || H <= 0 || F <= 0 || E <= 0 || k <= 0 || k > E) return 0;
    return dymoe::ffn_layout(T, H, F, E, k).total;
}

// Paper Sec. 4.3: cosine retention ratio, then the ceiling.  The product is
// lowered by 1e-9 before the ceiling so that an exactly integral r(l)*M that
// evaluates one ulp high (cos(pi/3) = 0.5000000000000001) is not rounded up.
int dymoe_depth_schedule(int layer, int n_layers, double lambda, int M)
{
    if (M < 1 || n_layers < 1 || layer < 0 || layer >= n_layers) return DYMOE_EINVAL;
    if (!(lambda >= 0.0 && lambda <= 1.0)) return DYMOE_EINVAL;
    double r = 1.0;
    if (n_layers > 1) {
        const double kPi = 3.141592653589793238462643383279502884;
        double c = cos(kPi * (double)layer / (double)(n_layers - 1));
        r = (1.0 - lambda) * 0.5 * (c + 1.0) + lambda;
    }
    double t = ceil(r * (double)M - 1e-9);
    if (t < 1.0) t = 1.0;
    if (t > (double)M) t = (double)M;
    return (int)t;
}

}  // extern "C"
