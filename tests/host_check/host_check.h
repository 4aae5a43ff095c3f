// Interface between the launcher stand-ins (stubs.cpp) and the driver of the host-side sanitizer test.
#ifndef HOST_CHECK_H_
#define HOST_CHECK_H_
#include <stddef.h>
#ifdef __cplusplus
extern "C" {
#endif
void hc_add_range(const void* p, size_t bytes, const char* name);   // memory a kernel may touch
void hc_clear_ranges(void);
void hc_set_mode(int mode);     // 0: tuned kernels refuse every shape, 1: they accept what the real ones would
long hc_checked(void);          // buffers checked so far
long hc_launches(void);         // launches seen so far
void* hc_scratch_address(void); // the address hipGetSymbolAddress reports for the static scratch array (driver's)
#ifdef __cplusplus
}
#endif
#endif
