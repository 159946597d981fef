#ifndef HIPMOCK_RUNTIME_H
#define HIPMOCK_RUNTIME_H
#include "hip_runtime_api.h"
#endif
