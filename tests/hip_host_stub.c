/* A stand-in for the HIP runtime, for host-only builds of the library under sanitizers
 * (tests/test_api_sanitizers.py): the handful of runtime entry points the library's host code refers
 * to.  Registration of device code does nothing; anything that would launch a kernel ends the
 * process, because the driver of that test must stay on the host side of every entry point. */
#include <stdio.h>
#include <stdlib.h>

static void no_launch(const char* what)
{
    fprintf(stderr, "host-only build: %s was reached (a kernel launch)\n", what);
    abort();
}

void** __hipRegisterFatBinary(const void* data) { static void* handle; (void)data; return &handle; }
void __hipUnregisterFatBinary(void** handle) { (void)handle; }
void __hipRegisterFunction(void** h, const void* f, char* a, const char* b, unsigned c, void* d, void* e, void* g, void* i, int* j)
{
    (void)h; (void)f; (void)a; (void)b; (void)c; (void)d; (void)e; (void)g; (void)i; (void)j;
}
void __hipRegisterVar(void** h, void* v, char* a, const char* b, int c, size_t d, int e, int g)
{
    (void)h; (void)v; (void)a; (void)b; (void)c; (void)d; (void)e; (void)g;
}
int __hipPushCallConfiguration(void) { no_launch("__hipPushCallConfiguration"); return 1; }
int __hipPopCallConfiguration(void) { no_launch("__hipPopCallConfiguration"); return 1; }
int hipLaunchKernel(void) { no_launch("hipLaunchKernel"); return 1; }
int hipGetLastError(void) { return 0; }
const char* hipGetErrorString(int e) { (void)e; return "no HIP runtime in this build"; }
int hipGetDevice(int* dev) { *dev = 0; return 0; }
int hipFuncSetAttribute(const void* f, int attr, int value) { (void)f; (void)attr; (void)value; return 0; }
int hipDeviceGetAttribute(int* value, int attr, int dev) { (void)attr; (void)dev; *value = 256; return 0; }
int hipGetSymbolAddress(void** p, const void* symbol) { (void)symbol; *p = NULL; return 1; }
