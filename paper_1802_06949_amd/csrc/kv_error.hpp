// Message behind kv_last_error(NULL): the last failure, on this thread, of a call that has no store.
#pragma once
void kv_set_global_error(const char* message);
