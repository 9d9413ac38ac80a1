// Kernels that need more dynamic LDS than the default limit announce it at load time, not at
// their first launch: instantiating a launcher odr-uses LdsAttr<kernel, bytes>::reg, whose
// constructor runs with the library's static initialisers and appends (kernel, bytes) to a list.
// No HIP call is made there.  The library's per-device set-up (see moc_api.hip) walks the list once
// per device and calls hipFuncSetAttribute for every entry, so no launcher keeps a "first call"
// flag and a first call may be made under stream capture.
#pragma once
#include <vector>

namespace moc {

struct KernelAttr {
    const void* fn;
    int lds_bytes;
};

inline std::vector<KernelAttr>& kernel_attr_list() {
    static std::vector<KernelAttr> v;
    return v;
}

template <auto Kern, int BYTES> struct LdsAttr {
    struct Reg {
        Reg() { kernel_attr_list().push_back(KernelAttr{reinterpret_cast<const void*>(Kern), BYTES}); }
    };
    static Reg reg;
    static inline void use() { (void)&reg; }
};
template <auto Kern, int BYTES> typename LdsAttr<Kern, BYTES>::Reg LdsAttr<Kern, BYTES>::reg;

constexpr int kMaxDynLds = 160 * 1024 - 64;   // what a workgroup may ask for on gfx950, minus the static use of the kernels here

}  // namespace moc
