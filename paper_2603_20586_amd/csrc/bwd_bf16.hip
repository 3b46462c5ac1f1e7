// placeholder, replaced below
#include "mka_dev.h"
#include "mka_internal.h"
namespace mka {
size_t bwd_workspace_bytes(int BH, int Tq, int S, int d) { (void)BH; (void)Tq; (void)S; (void)d; return 256; }
hipError_t launch_bwd_bf16(const BwdArgs& a, hipStream_t st) { (void)a; (void)st; return hipErrorNotSupported; }
}
