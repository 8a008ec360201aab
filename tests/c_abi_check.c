/* Plain C99 user of include/soar.h: the header compiles as C, every entry point links, the
 * structure layouts are the ones the Python binding assumes (sizes and offsets are printed for the
 * test to compare), and host-side validation answers without a GPU.  Built and run by
 * tests/test_abi.py; no compute call is made. */
#include <stddef.h>
#include <stdio.h>
#include <string.h>

#include "soar.h"

#define SHOW(type, field) printf(#type "." #field " %zu\n", offsetof(type, field))

int main(void)
{
    soar_params p;
    soar_mx_params mp;
    soar_tensor_desc d;
    typedef void (*any_fn)(void);
    any_fn fns[] = {
        (any_fn)soar_default_params, (any_fn)soar_paper_params, (any_fn)soar_workspace_bytes,
        (any_fn)soar_quantize, (any_fn)soar_quantize_static, (any_fn)soar_quantize_batch, (any_fn)soar_batch_workspace_bytes,
        (any_fn)soar_dequantize, (any_fn)soar_recon_error, (any_fn)soar_dequantize_batch,
        (any_fn)soar_recon_error_batch, (any_fn)soar_e2m1_round_f32, (any_fn)soar_e4m3_project_f32,
        (any_fn)soar_rcp_midrange_f32, (any_fn)soar_mx_default_params, (any_fn)soar_mxfp4_workspace_bytes,
        (any_fn)soar_mxfp4_quantize, (any_fn)soar_mxfp4_quantize_batch, (any_fn)soar_mxfp4_batch_workspace_bytes,
        (any_fn)soar_mxfp4_dequantize, (any_fn)soar_mxfp4_dequantize_batch, (any_fn)soar_kernel_timing_enable, (any_fn)soar_kernel_timing_read, (any_fn)soar_search_stats_enable, (any_fn)soar_search_stats_read, (any_fn)soar_debug_arrival_plan,
        (any_fn)soar_status_string, (any_fn)soar_version,
    };
    size_t k;
    for (k = 0; k < sizeof(fns) / sizeof(fns[0]); ++k)
        if (!fns[k]) return 1;

    printf("sizeof soar_params %zu\n", sizeof(soar_params));
    printf("sizeof soar_tensor_desc %zu\n", sizeof(soar_tensor_desc));
    printf("sizeof soar_stored_desc %zu\n", sizeof(soar_stored_desc));
    printf("sizeof soar_mx_params %zu\n", sizeof(soar_mx_params));
    printf("sizeof soar_mx_tensor_desc %zu\n", sizeof(soar_mx_tensor_desc));
    SHOW(soar_params, dss_radius);
    SHOW(soar_params, early_stop_rel);
    SHOW(soar_params, streams);
    SHOW(soar_tensor_desc, d_codes);
    SHOW(soar_tensor_desc, d_amax_in);
    SHOW(soar_stored_desc, dtype);
    SHOW(soar_stored_desc, d_sse);
    SHOW(soar_mx_params, radius);
    SHOW(soar_mx_params, streams);
    SHOW(soar_mx_tensor_desc, d_status);

    soar_default_params(&p);
    soar_mx_default_params(&mp);
    printf("default iters %d n_beta %d block %d struct_size %u\n", (int)p.iters, (int)p.n_beta, (int)p.block,
           (unsigned)p.struct_size);
    printf("version %u\n", (unsigned)soar_version());
    printf("workspace 256x256 %zu\n", soar_workspace_bytes(256, 256, &p));
    printf("null weights %d\n", (int)soar_quantize(NULL, SOAR_BF16, 4, 64, 64, &p, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL));
    memset(&d, 0, sizeof(d));
    printf("empty batch %d\n", (int)soar_quantize_batch(0, &d, &p, NULL, 0, NULL));
    printf("bad shape %d\n", (int)soar_dequantize((const uint8_t *)8, (const uint8_t *)16, (const float *)32, 4, 60,
                                                  SOAR_BF16, (void *)4096, 64, NULL));
    printf("status text %s\n", soar_status_string(SOAR_ERR_SHAPE));
    return 0;
}
