// Declarations shared by the library's own translation units (not part of the C boundary).
#ifndef PSGD_INTERNAL_H
#define PSGD_INTERNAL_H

namespace psgd {

// Records a printf-style message for psgd_last_error() on this thread and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

}  // namespace psgd

#endif
