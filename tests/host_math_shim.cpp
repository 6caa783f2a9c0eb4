// Host build of the library's noise arithmetic (the same header the kernels include), so that its
// logic can be checked on a machine without a GPU.  Not part of the product.
#include "../paper_2507_01154_amd/csrc/philox_gauss.h"
extern "C" {
void shim_philox(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
  flashdp::Words4 w = flashdp::philox4x32_10(ctr[0], ctr[1], ctr[2], ctr[3], key[0], key[1]);
  for (int i = 0; i < 4; ++i) out[i] = w.w[i];
}
void shim_box_muller(const uint32_t* words, long n_groups, float* z) {
  for (long g = 0; g < n_groups; ++g) {
    flashdp::Words4 w;
    for (int i = 0; i < 4; ++i) w.w[i] = words[4 * g + i];
    flashdp::Normals4 o = flashdp::box_muller4(w);
    for (int i = 0; i < 4; ++i) z[4 * g + i] = o.z[i];
  }
}
void shim_noise_field(uint64_t seed, uint32_t layer, long n, float* z) {
  for (long g = 0; 4 * g < n; ++g) {
    flashdp::Normals4 o = flashdp::noise_group(seed, layer, (uint64_t)g);
    for (int i = 0; i < 4 && 4 * g + i < n; ++i) z[4 * g + i] = o.z[i];
  }
}
}
