/*
 * wap_testing.h -- hooks of libwap that exist for its parity tests only; not part of the product boundary.
 */
#ifndef WAP_TESTING_H
#define WAP_TESTING_H

#ifdef __cplusplus
extern "C" {
#endif

/* Process-wide and NOT thread safe (plain globals read while a plan is made): force the tile configuration of
 * the forward-type kernels (0..9), of the weight-gradient kernel (0..4; 5 / 6: the patch kernel with two / one
 * 32-channel dy blocks per wavefront) and the number of reduction splits;
 * -1 restores the shape-driven choice.  Forced values that the shape cannot use are ignored, and the
 * *_workspace_bytes queries reflect the forced choice.  Lets the tests reach every kernel and tile
 * configuration with small shapes. */
void wap_debug_force(int fwd_cfg, int wgrad_cfg, int nsplit);

#ifdef __cplusplus
}
#endif
#endif /* WAP_TESTING_H */
