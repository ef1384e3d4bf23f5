// Host-only driver for the sanitizer build of the planner (address + undefined behaviour): plans layer shapes read from
// stdin (nine integers per line: N C H W K R S pad_h pad_w) with every host-only entry point, then requests every tile
// shape of every family with every loader, every work-group numbering and a few share counts. Touches no device. Prints the number of plans made.
#include "../../include/convfwd.h"

#include <cstdio>
#include <cstring>

int main()
{
    int d[9];
    long plans = 0, refused = 0;
    while (std::scanf("%d %d %d %d %d %d %d %d %d", &d[0], &d[1], &d[2], &d[3], &d[4], &d[5], &d[6], &d[7], &d[8]) == 9) {
        conv_plan_t p, q;
        const int rc = conv_fwd_plan(d[0], d[1], d[2], d[3], d[4], d[5], d[6], d[7], d[8], &p);
        if (rc != CONV_OK) { ++refused; continue; }
        ++plans;
        if (conv_fwd_plan_split_c(d[0], d[1], d[2], d[3], d[4], d[5], d[6], d[7], d[8], &q) == CONV_OK) ++plans;
        (void)conv_two_stage_workspace_bytes(d[0], d[1], d[2], d[3], d[4], d[5], d[6], d[7], d[8]);
        for (int kernel = 0; kernel <= 3; ++kernel) {
            const int nv = conv_variant_count(kernel);
            for (int v = 0; v < nv; ++v) {
                for (int loader = 0; loader <= 4; ++loader) {
                    for (int shares = 0; shares <= 5; shares += 5) {
                        conv_plan_t req;
                        std::memset(&req, 0, sizeof(req));
                        req.kernel = kernel; req.variant = v; req.loader = loader; req.c_splits = shares;
                        req.order = (v + shares) % 4; req.k_group = req.order == 3 ? (v % 3) * 2 : 0;
                        req.tile_pix = (v + loader) % 3 == 0 ? 0 : 1 + (v * 37 + loader * 11) % 97;
                        double cycles = 0;
                        const int r2 = conv_fwd_plan_request(d[0], d[1], d[2], d[3], d[4], d[5], d[6], d[7], d[8], &req, &q, &cycles);
                        if (r2 == CONV_OK) ++plans; else ++refused;
                        if (kernel != CONV_KERNEL_TAP) break;
                    }
                    if (kernel != CONV_KERNEL_TAP) break;
                }
            }
        }
    }
    for (int code = 1; code >= -9; --code) (void)conv_strerror(code);
    std::printf("plans %ld refused %ld\n", plans, refused);
    return plans > 0 ? 0 : 1;
}
